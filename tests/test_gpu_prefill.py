"""GPU parity of jd_prefill_attention (causal attention of new tokens over the paged cache) against the fp64
oracle, element by element, to the decode path's tolerance (max-abs 5e-3, max-rel 1e-2 above the floor)."""
import numpy as np
import pytest

from paper_2604_23838_amd import workloads as W
from helpers import error_report, prefill_inputs

pytestmark = pytest.mark.gpu

ABS_TOL, REL_TOL = 5e-3, 1e-2


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    return torch


def bf16_dev(torch, a):
    return torch.from_numpy(a.view(np.int16)).to("cuda:0").view(torch.bfloat16)


def run_prefill(torch, w, q, q_lens, offs, max_q_len=None, scale=0.0):
    from paper_2604_23838_amd import binding as jb
    s = w.shape
    op = jb.DecodeAttention(s.batch, s.num_q_heads, s.num_kv_heads, s.head_dim, w.max_pages_per_seq, w.num_pages,
                            softmax_scale=scale)
    out = torch.full(q.shape, 777.0, dtype=torch.float32, device="cuda:0")     # sentinel: unowned rows stay put
    op.prefill(bf16_dev(torch, q), bf16_dev(torch, w.k_pages), bf16_dev(torch, w.v_pages),
               torch.from_numpy(w.block_table).to("cuda:0"), torch.from_numpy(w.seq_lens).to("cuda:0"),
               torch.from_numpy(np.asarray(q_lens, dtype=np.int32)).to("cuda:0"),
               torch.from_numpy(np.asarray(offs, dtype=np.int32)).to("cuda:0"),
               int(max(q_lens)) if max_q_len is None else max_q_len, out=out)
    torch.cuda.synchronize()
    op.check_flags()
    op.close()
    return out.cpu().numpy()


def check(got, ref, q_lens, offs):
    owned = np.zeros(got.shape[0], dtype=bool)
    for b, n in enumerate(q_lens):
        owned[offs[b]:offs[b] + n] = True
    assert np.all(got[~owned] == 777.0), "rows of no request were written"
    if owned.any():
        assert np.isfinite(got[owned]).all()
        ma, mr = error_report(got[owned], ref[owned])
        assert ma <= ABS_TOL and mr <= REL_TOL, (ma, mr)


SHAPES = [(8, 2, 64), (32, 8, 128), (14, 2, 64), (64, 8, 128), (16, 1, 64), (12, 4, 128), (4, 4, 128), (16, 16, 64), (48, 24, 128)]


@pytest.mark.parametrize("hq,hkv,d", SHAPES)
def test_chunks_after_a_context_and_full_prefills(torch_cuda, jo, hq, hkv, d):
    shp = W.Shape("t", 0, hq, hkv, d, 1)
    lens = np.array([17, 100, 250, 1000, 16, 1, 333, 48, 5], dtype=np.int32)
    # full prefill, chunk after a context, nothing to do, one token (= decode), ragged tails, page-aligned
    ql = np.array([17, 33, 0, 257, 16, 1, 1, 32, 3], dtype=np.int32)
    w = W.build(shp, lens, seed=5, cfg=81)
    q, ql, offs = prefill_inputs(w, ql, seed=6)
    ref = jo.prefill_attention(q, w.k_pages, w.v_pages, w.block_table, w.seq_lens, ql, offs)
    got = run_prefill(torch_cuda, w, q, ql, offs)
    check(got, ref, ql, offs)


def test_single_new_token_equals_the_decode_entry_point(torch_cuda, jo):
    from paper_2604_23838_amd import binding as jb
    torch = torch_cuda
    w = W.gen_config(1, 3)
    s = w.shape
    ql = np.ones(s.batch, dtype=np.int32)
    offs = np.arange(s.batch, dtype=np.int32)
    got = run_prefill(torch, w, w.q, ql, offs)
    op = jb.DecodeAttention(s.batch, s.num_q_heads, s.num_kv_heads, s.head_dim, w.max_pages_per_seq, w.num_pages)
    dec = op(bf16_dev(torch, w.q), bf16_dev(torch, w.k_pages), bf16_dev(torch, w.v_pages),
             torch.from_numpy(w.block_table).to("cuda:0"), torch.from_numpy(w.seq_lens).to("cuda:0"))
    torch.cuda.synchronize()
    ref = jo.decode_attention(w.q, w.k_pages, w.v_pages, w.block_table, w.seq_lens)
    check(got, ref, ql, offs)
    assert np.abs(got - dec.cpu().numpy()).max() <= 1e-5


def _set_keys_along(w, b, direction, gain):
    """Keys of request b become gain[t] * direction at position t (every kv head), through the block table."""
    for t in range(int(w.seq_lens[b])):
        page, slot = int(w.block_table[b, t // 16]), t % 16
        w.k_pages[page, :, slot, :] = W.f32_to_bf16_bits((gain[t] * direction).astype(np.float32))


@pytest.mark.parametrize("hq,hkv,d", [(32, 8, 128), (14, 2, 64)])
def test_scores_that_outgrow_the_reference_exponent(torch_cuda, jo, hq, hkv, d):
    """The kernel keeps a row's reference exponent until the row's probabilities outgrow it.  Scores that climb
    along the sequence by several binades a token force that re-centring tile after tile; a single spike in
    mid-sequence forces it once, by 100 binades; falling scores never do.  Every row against the oracle."""
    shp = W.Shape("t", 0, hq, hkv, d, 1)
    lens = np.array([700, 431, 520, 300], dtype=np.int32)
    ql = np.array([700, 200, 520, 300], dtype=np.int32)
    w = W.build(shp, lens, seed=21, cfg=86)
    q, ql, offs = prefill_inputs(w, ql, seed=22)
    u = np.zeros(d, dtype=np.float64)
    u[: d // 2] = 1.0                                   # |u|^2 = d / 2, so q . k = gain * d / 2 for q = u
    per_unit = (d / 2) / np.sqrt(d) * np.log2(np.e)     # binades of score per unit of gain
    ramps = [np.arange(700) * (2.5 / per_unit),          # +2.5 binades a token: 80 a tile
             np.where(np.arange(431) == 300, 100.0 / per_unit, 0.0),   # one key 100 binades above the rest
             -np.arange(520) * (1.0 / per_unit),         # falling: the first tile's reference stays
             np.sin(np.arange(300) * 0.05) * (40.0 / per_unit)]        # rising and falling by 40 binades
    for b, g in enumerate(ramps):
        _set_keys_along(w, b, u, g)
        q[offs[b]:offs[b] + ql[b]] = W.f32_to_bf16_bits(np.broadcast_to(u, (int(ql[b]), hq, d)).astype(np.float32))
    ref = jo.prefill_attention(q, w.k_pages, w.v_pages, w.block_table, w.seq_lens, ql, offs)
    got = run_prefill(torch_cuda, w, q, ql, offs)
    check(got, ref, ql, offs)


def test_long_prefill_spans_many_query_blocks(torch_cuda, jo):
    shp = W.Shape("t", 0, 32, 8, 128, 1)
    lens = np.array([3000, 1111, 4097], dtype=np.int32)
    ql = np.array([3000, 600, 1025], dtype=np.int32)
    w = W.build(shp, lens, seed=9, cfg=82)
    q, ql, offs = prefill_inputs(w, ql, seed=10)
    ref = jo.prefill_attention(q, w.k_pages, w.v_pages, w.block_table, w.seq_lens, ql, offs)
    got = run_prefill(torch_cuda, w, q, ql, offs)
    check(got, ref, ql, offs)


def test_scale_override_and_bound_on_query_length(torch_cuda, jo):
    shp = W.Shape("t", 0, 8, 2, 64, 1)
    lens = np.array([200, 90], dtype=np.int32)
    ql = np.array([120, 90], dtype=np.int32)
    w = W.build(shp, lens, seed=11, cfg=83)
    q, ql, offs = prefill_inputs(w, ql, seed=12)
    ref = jo.prefill_attention(q, w.k_pages, w.v_pages, w.block_table, w.seq_lens, ql, offs, scale=0.2)
    got = run_prefill(torch_cuda, w, q, ql, offs, max_q_len=4096, scale=0.2)     # a loose bound is fine
    check(got, ref, ql, offs)


def test_no_new_tokens_writes_nothing(torch_cuda, jo):
    shp = W.Shape("t", 0, 8, 2, 64, 1)
    w = W.build(shp, np.array([40, 0, 7], dtype=np.int32), seed=13, cfg=84)
    q, ql, offs = prefill_inputs(w, [0, 0, 0], seed=14)
    got = run_prefill(torch_cuda, w, q, ql, offs, max_q_len=0)
    assert np.all(got == 777.0)
    got = run_prefill(torch_cuda, w, q, ql, offs, max_q_len=64)
    assert np.all(got == 777.0)


def test_bad_page_id_is_flagged_not_dereferenced(torch_cuda):
    from paper_2604_23838_amd import binding as jb
    w = W.gen_config(1, 0)
    bt = w.block_table.copy()
    bt[3, 40] = w.num_pages + 12345       # a page in the middle of the longest request
    bt[1, 0] = -7
    bad = W.Workload(w.cfg, w.seed, w.shape, w.q, w.k_pages, w.v_pages, bt, w.seq_lens)
    ql = np.array([5, 100, 0, 64], dtype=np.int32)
    q, ql, offs = prefill_inputs(bad, ql, seed=3)
    with pytest.raises(jb.JdError) as e:
        run_prefill(torch_cuda, bad, q, ql, offs)
    assert e.value.status == jb.JD_ERR_BAD_INPUT


def test_random_shapes_and_chunks(torch_cuda, jo):
    # a seeded sweep over head layouts, both head sizes, contexts and chunk lengths
    rng = np.random.default_rng(77)
    heads = [(1, 1), (3, 1), (5, 5), (6, 2), (8, 8), (12, 4), (16, 2), (16, 1), (24, 8), (40, 8)]
    for case in range(16):
        hq, hkv = heads[rng.integers(len(heads))]
        d = int(rng.choice([64, 128]))
        B = int(rng.integers(1, 12))
        lens = np.floor(rng.lognormal(np.log(200.0), 1.2, size=B)).clip(0, 3000).astype(np.int32)
        frac = rng.random(B)
        ql = np.where(rng.random(B) < 0.25, lens, np.floor(lens * frac)).astype(np.int32)   # whole prompts and chunks
        ql = np.minimum(ql, 700)
        w = W.build(W.Shape("t", 0, hq, hkv, d, 1), lens, seed=100 + case, cfg=85)
        q, ql, offs = prefill_inputs(w, ql, seed=200 + case)
        ref = jo.prefill_attention(q, w.k_pages, w.v_pages, w.block_table, w.seq_lens, ql, offs)
        got = run_prefill(torch_cuda, w, q, ql, offs, max_q_len=int(max(int(ql.max()), 1)))
        check(got, ref, ql, offs)


def test_repeated_calls_are_bitwise_identical(torch_cuda):
    # nothing in the kernel depends on timing: the same inputs give the same bits, call after call
    shp = W.Shape("t", 0, 10, 2, 128, 1)
    lens = np.array([1500, 77, 1030, 2600, 640], dtype=np.int32)
    ql = np.array([1500, 22, 700, 300, 640], dtype=np.int32)
    w = W.build(shp, lens, seed=31, cfg=87)
    q, ql, offs = prefill_inputs(w, ql, seed=32)
    first = run_prefill(torch_cuda, w, q, ql, offs)
    for _ in range(4):
        again = run_prefill(torch_cuda, w, q, ql, offs)
        assert np.array_equal(first.view(np.uint32), again.view(np.uint32))


def test_wide_batch_of_tiny_chunks(torch_cuda, jo):
    # thousands of requests with zero to a few new tokens each: the ranking kernel runs over many tiles and
    # most blocks of the launch have a single, mostly padded, tile of rows
    rng = np.random.default_rng(61)
    B = 2500
    lens = rng.integers(0, 90, size=B).astype(np.int32)
    ql = np.minimum(lens, rng.integers(0, 4, size=B)).astype(np.int32)
    w = W.build(W.Shape("t", 0, 14, 2, 64, 1), lens, seed=61, cfg=86)
    q, ql, offs = prefill_inputs(w, ql, seed=62)
    ref = jo.prefill_attention(q, w.k_pages, w.v_pages, w.block_table, w.seq_lens, ql, offs)
    got = run_prefill(torch_cuda, w, q, ql, offs, max_q_len=3)
    check(got, ref, ql, offs)


def test_hip_graph_capture_and_replay(torch_cuda, jo):
    # the call only enqueues two kernels: it can be captured, and every replay (eager work and synchronisations in
    # between, new chunk lengths written into the captured buffers) must match the oracle
    from paper_2604_23838_amd import binding as jb
    torch = torch_cuda
    shp = W.Shape("t", 0, 12, 4, 128, 1)
    lens = np.array([900, 130, 2049, 64, 555], dtype=np.int32)
    w = W.build(shp, lens, seed=41, cfg=88)
    cap = 600                                     # the captured launch is sized for chunks of up to 600 tokens
    q, _, _ = prefill_inputs(w, np.full(len(lens), cap, dtype=np.int32), seed=42)
    offs = (np.arange(len(lens)) * cap).astype(np.int32)
    op = jb.DecodeAttention(len(lens), shp.num_q_heads, shp.num_kv_heads, shp.head_dim, w.max_pages_per_seq, w.num_pages)
    tq, tk, tv = bf16_dev(torch, q), bf16_dev(torch, w.k_pages), bf16_dev(torch, w.v_pages)
    tbt, tl = torch.from_numpy(w.block_table).to("cuda:0"), torch.from_numpy(w.seq_lens).to("cuda:0")
    ql = np.minimum(lens, [600, 100, 300, 64, 1]).astype(np.int32)
    tql, tof = torch.from_numpy(ql).to("cuda:0"), torch.from_numpy(offs).to("cuda:0")
    out = torch.full(q.shape, 777.0, dtype=torch.float32, device="cuda:0")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        op.prefill(tq, tk, tv, tbt, tl, tql, tof, cap, out=out)      # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    eager = out.cpu().numpy().copy()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        op.prefill(tq, tk, tv, tbt, tl, tql, tof, cap, out=out)
    rng = np.random.default_rng(5)
    for rep in range(4):
        if rep:
            ql = np.minimum(lens, rng.integers(0, cap + 1, size=len(lens))).astype(np.int32)
            tql.copy_(torch.from_numpy(ql))
        out.fill_(777.0)                          # eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        ref = jo.prefill_attention(q, w.k_pages, w.v_pages, w.block_table, w.seq_lens, ql, offs)
        check(got, ref, ql, offs)
        if rep == 0:
            assert np.array_equal(got.view(np.uint32), eager.view(np.uint32))
    op.check_flags()
    op.close()


def sampled_token_check(torch_cuda, jo, w, q, ql, offs, got, per_request=3, seed=3):
    """Token t of request b's new tokens is the decode step of its first c + t + 1 tokens (c = context): pinned
    on the CPU (a one-token prefill is bitwise the decode oracle, later tokens never influence earlier ones)."""
    pick = np.random.default_rng(seed)
    samples = []
    for b in range(len(ql)):
        n = int(ql[b])
        if n == 0:
            continue
        fixed = [0, 1, 15, 16, 31, 32, 63, 64, 127, 128, n // 2, n - 65, n - 2, n - 1]
        for t in fixed[:4] + fixed[-4:] if b % 4 else fixed:
            samples.append((b, min(max(t, 0), n - 1)))
        for t in pick.integers(0, n, size=per_request):
            samples.append((b, int(t)))
    sb = np.array([s_[0] for s_ in samples]); st = np.array([s_[1] for s_ in samples])
    ctx = (w.seq_lens.astype(np.int64) - ql)[sb]
    q_dec = np.ascontiguousarray(q[offs[sb] + st])                      # [S, Hq, D]
    bt_dec = np.ascontiguousarray(w.block_table[sb])
    len_dec = (ctx + st + 1).astype(np.int32)
    ref = jo.decode_attention(q_dec, w.k_pages, w.v_pages, bt_dec, len_dec)
    g = got[offs[sb] + st]
    assert np.isfinite(g).all()
    ma, mr = error_report(g, ref)
    print(f"{len(samples)} sampled tokens: max-abs {ma:.3e} max-rel {mr:.3e}", flush=True)
    assert ma <= ABS_TOL and mr <= REL_TOL, (ma, mr)


@pytest.mark.parametrize("cfg,new_turn", [(2, 0), (4, 0), (5, 0), (2, 512), (4, 512), (5, 512)])
def test_full_size_on_sampled_tokens(torch_cuda, jo, cfg, new_turn):
    # The benchmark's prefill workloads at full size on the three benchmark head shapes (G = 4; G = 8; head_dim 64
    # with G = 7): the first 32 requests of the config's length draw, recomputed whole (new_turn = 0: what a
    # migrated request costs its target) or as the context of a new 512-token turn.  The whole oracle output would
    # take hours, so sampled tokens are checked one by one.
    lens = W.draw_seq_lens(cfg, np.random.default_rng(0))[:32].astype(np.int32)
    shp = W.SHAPES[cfg]
    w = W.build(W.Shape("p", 0, shp.num_q_heads, shp.num_kv_heads, shp.head_dim, 1), lens + new_turn, seed=1, cfg=70,
                threads=16)
    ql = np.full(len(lens), new_turn, dtype=np.int32) if new_turn else lens.copy()
    q, ql, offs = prefill_inputs(w, ql, seed=2)
    got = run_prefill(torch_cuda, w, q, ql, offs)
    sampled_token_check(torch_cuda, jo, w, q, ql, offs, got)


def test_prefill_and_decode_alternate_on_one_handle(torch_cuda, jo):
    # one handle, one stream: prefill of new turns, a decode step, another prefill with other lengths, another
    # decode step; the two calls share the handle's workspace and must leave nothing behind for each other
    from paper_2604_23838_amd import binding as jb
    torch = torch_cuda
    shp = W.SHAPES[5]
    lens = np.array([700, 33, 0, 5000, 260, 16, 2049, 1], dtype=np.int32)
    w = W.build(shp, lens, seed=8, cfg=96)
    B = len(lens)
    tk, tv = bf16_dev(torch, w.k_pages), bf16_dev(torch, w.v_pages)
    tbt, tl = torch.from_numpy(w.block_table).to("cuda:0"), torch.from_numpy(lens).to("cuda:0")
    tqd = bf16_dev(torch, w.q)
    op = jb.DecodeAttention(B, shp.num_q_heads, shp.num_kv_heads, shp.head_dim, w.max_pages_per_seq, w.num_pages)
    rng = np.random.default_rng(9)
    for step in range(3):
        cur = lens if step == 0 else np.minimum(lens, rng.integers(0, 5001, size=B)).astype(np.int32)
        tl.copy_(torch.from_numpy(cur))
        ql = np.minimum(cur, rng.integers(0, 400, size=B)).astype(np.int32)
        q, ql, offs = prefill_inputs(w, ql, seed=10 + step)
        outp = torch.full(q.shape, 777.0, dtype=torch.float32, device="cuda:0")
        op.prefill(bf16_dev(torch, q), tk, tv, tbt, tl, torch.from_numpy(ql).to("cuda:0"),
                   torch.from_numpy(offs[:B].astype(np.int32)).to("cuda:0"), int(max(int(ql.max()), 1)), out=outp)
        outd = torch.full((B, shp.num_q_heads, shp.head_dim), float("nan"), dtype=torch.float32, device="cuda:0")
        op(tqd, tk, tv, tbt, tl, outd)
        torch.cuda.synchronize()
        check(outp.cpu().numpy(), jo.prefill_attention(q, w.k_pages, w.v_pages, w.block_table, cur, ql, offs), ql, offs)
        refd = jo.decode_attention(w.q, w.k_pages, w.v_pages, w.block_table, cur)
        gd = outd.cpu().numpy()
        assert np.isfinite(gd).all()
        ma, mr = error_report(gd, refd)
        assert ma <= ABS_TOL and mr <= REL_TOL, (step, ma, mr)
    op.check_flags()
    op.close()


def test_query_rows_outside_the_buffers_are_skipped_and_flagged(torch_cuda, jo):
    # a request whose offset and length leave [0, TQ) is not computed at all (nothing of it is read or written)
    # and raises the sticky flag; its neighbours are unaffected
    from paper_2604_23838_amd import binding as jb
    torch = torch_cuda
    w = W.gen_config(1, 0)
    ql = np.array([5, 20, 0, 64], dtype=np.int32)
    q, ql, offs = prefill_inputs(w, ql, seed=4)
    TQ = q.shape[0]
    s = w.shape
    for bad_off in (TQ - 10, -3):
        o2 = offs[:4].astype(np.int32).copy()
        o2[1] = bad_off                         # request 1 (20 new tokens) would run past the end / start before 0
        op = jb.DecodeAttention(s.batch, s.num_q_heads, s.num_kv_heads, s.head_dim, w.max_pages_per_seq, w.num_pages)
        out = torch.full(q.shape, 777.0, dtype=torch.float32, device="cuda:0")
        op.prefill(bf16_dev(torch, q), bf16_dev(torch, w.k_pages), bf16_dev(torch, w.v_pages),
                   torch.from_numpy(w.block_table).to("cuda:0"), torch.from_numpy(w.seq_lens).to("cuda:0"),
                   torch.from_numpy(ql).to("cuda:0"), torch.from_numpy(o2).to("cuda:0"), 64, out=out)
        torch.cuda.synchronize()
        with pytest.raises(jb.JdError) as e:
            op.check_flags()
        assert e.value.status == jb.JD_ERR_BAD_INPUT and "query rows" in str(e.value)
        op.close()
        got = out.cpu().numpy()
        ql_ok = ql.copy(); ql_ok[1] = 0
        ref = jo.prefill_attention(q, w.k_pages, w.v_pages, w.block_table, w.seq_lens, ql_ok, offs)
        check(got, ref, ql_ok, offs)            # request 1's rows still hold the sentinel, the others are right
