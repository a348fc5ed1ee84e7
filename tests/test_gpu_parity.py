"""GPU parity: libjigsaw_decode (through the C ABI binding) against the fp64 CPU oracle.

Tolerance (stated by the benchmark spec): max-abs <= 5e-3 and max-rel <= 1e-2, both required, where
max-rel is |g - o| / max(|o|, 1e-3) (outputs of diffuse softmax over N(0,1) values are ~1e-2
in magnitude and cross zero, so an un-floored element-wise ratio would only measure fp32
rounding noise).  The kernels accumulate in fp32 and land around 1e-6, far inside both.
"""
import numpy as np
import pytest

from paper_2604_23838_amd import workloads as W
from gpu_helpers import arrays, check, run_gpu, to_dev
from helpers import pack_paged

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (run with -m 'not gpu' elsewhere)")
    return torch


def test_tiny_config(torch_cuda, jo):
    w = W.gen_config(1, 0)
    ref = jo.decode_attention(*arrays(w))
    check(run_gpu(torch_cuda, arrays(w)), ref, f"cfg1")


EDGE_LENS = [
    [1], [15], [16], [17], [31, 32, 33], [0, 5, 0], [0, 0, 0], [1, 1, 1, 1, 1, 1, 1, 1, 1],
    [1000, 1, 0, 64, 65], [4096], [63, 0, 0, 0, 0, 0, 0, 2049],
]


@pytest.mark.parametrize("shape", [(8, 2, 64), (14, 2, 64), (32, 8, 128), (64, 8, 128), (4, 4, 128), (16, 1, 64)])
def test_edge_lengths(torch_cuda, jo, shape):
    Hq, Hkv, D = shape
    for i, lens in enumerate(EDGE_LENS):
        rng = np.random.default_rng(1000 + i)
        q = rng.standard_normal((len(lens), Hq, D), dtype=np.float32)
        ks = [rng.standard_normal((L, Hkv, D), dtype=np.float32) for L in lens]
        vs = [rng.standard_normal((L, Hkv, D), dtype=np.float32) for L in lens]
        arrs = pack_paged(q, ks, vs, seed=i)
        ref = jo.decode_attention(*arrs)
        check(run_gpu(torch_cuda, arrs), ref, f"edge {lens} {shape}")


def test_ragged_batch_many_tiles(torch_cuda, jo):
    # long-tailed lengths spanning many spans, with a ragged tail on every request
    rng = np.random.default_rng(7)
    lens = np.clip(np.floor(rng.lognormal(np.log(600.0), 1.3, size=96)), 1, 20000).astype(np.int32)
    lens[5] = 0
    for shp in (W.SHAPES[2], W.SHAPES[5]):
        w = W.build(shp, lens, seed=7, cfg=90)
        ref = jo.decode_attention(*arrays(w))
        check(run_gpu(torch_cuda, arrays(w)), ref, f"ragged {shp.name}")


def test_wide_batch_of_short_requests(torch_cuda, jo):
    # more requests than threads in a block (the partition scan takes several requests per thread), many of
    # them empty or a single token
    rng = np.random.default_rng(12)
    lens = rng.integers(0, 70, size=3001).astype(np.int32)
    lens[rng.integers(0, 3001, size=600)] = 0
    lens[-1] = 777
    w = W.build(W.SHAPES[5], lens, seed=12, cfg=94)
    ref = jo.decode_attention(*arrays(w))
    check(run_gpu(torch_cuda, arrays(w)), ref, f"wide batch")


def test_one_very_long_sequence_cut_into_many_pieces(torch_cuda, jo):
    # 131 071 tokens in one request: each of its kv heads is cut over about a hundred waves, so the merge of the
    # pieces runs over several batches of records; the short neighbour shares the first wave with it
    lens = np.array([131071, 40], dtype=np.int32)
    w = W.build(W.SHAPES[2], lens, seed=23, cfg=91)
    ref = jo.decode_attention(*arrays(w))
    check(run_gpu(torch_cuda, arrays(w)), ref, f"very long")


@pytest.mark.parametrize("hq,hkv,d", [(14, 2, 64), (64, 4, 128), (8, 8, 128), (6, 6, 64), (16, 1, 128), (16, 1, 64), (24, 2, 64)])
def test_long_sequences_on_every_record_size(torch_cuda, jo, hq, hkv, d):
    # the merge of many pieces with 1, 2 and 4 KiB query slots (its batch size depends on it), group sizes 1 to 16,
    # wave groups of 1, 2 and 4, and every instantiation of the kernel (64-wide heads with a 2 KiB slot included)
    lens = np.array([7, 50000, 0, 33000], dtype=np.int32)
    w = W.build(W.Shape("t", 0, hq, hkv, d, 1), lens, seed=24, cfg=90)
    ref = jo.decode_attention(*arrays(w))
    check(run_gpu(torch_cuda, arrays(w)), ref, f"long sequences {hq}/{hkv}/{d}")


def test_largest_supported_batch(torch_cuda, jo):
    # the fused kernel keeps its partition tables in LDS, which bounds the batch at 8192 rows: all of them
    # live here, short, ragged, with a few long ones in between; one row more is refused at creation
    from paper_2604_23838_amd import binding as jb
    rng = np.random.default_rng(21)
    lens = rng.integers(1, 40, size=8192).astype(np.int32)
    lens[[5, 4000, 8191]] = [3000, 1500, 2049]
    w = W.build(W.SHAPES[5], lens, seed=21, cfg=92)
    ref = jo.decode_attention(*arrays(w))
    check(run_gpu(torch_cuda, arrays(w)), ref, "largest batch")
    s = W.SHAPES[5]
    cfg = jb.jd_config(8193, s.num_q_heads, s.num_kv_heads, s.head_dim, 16, 4, 64, 0.0, 0)
    with pytest.raises(jb.JdError) as e:
        jb.jd_create(cfg)
    assert e.value.status == jb.JD_ERR_UNSUPPORTED


def test_stragglers_scattered_in_a_finished_batch(torch_cuda, jo):
    # a big batch in which all but a few requests have finished: the walk from one live request to the next
    # crosses long runs of empty rows
    lens = np.zeros(3000, dtype=np.int32)
    lens[[0, 1, 70, 1029, 1030, 2998]] = [5000, 33, 7000, 16, 4097, 9000]
    w = W.build(W.SHAPES[2], lens, seed=13, cfg=99)
    ref = jo.decode_attention(*arrays(w))
    check(run_gpu(torch_cuda, arrays(w)), ref, f"scattered stragglers")


def test_scale_override_and_sharp_softmax(torch_cuda, jo):
    # large scale: the softmax is dominated by a few tokens; exercises the running-max rescale
    w = W.gen_config(1, 3)
    ref = jo.decode_attention(*arrays(w), scale=1.5)
    check(run_gpu(torch_cuda, arrays(w), scale=1.5), ref, f"scale 1.5")


def test_closed_forms_on_gpu(torch_cuda):
    # single key returns V exactly; zero query gives the mean over exactly L tokens
    rng = np.random.default_rng(21)
    q = rng.standard_normal((2, 8, 128), dtype=np.float32)
    ks = [rng.standard_normal((1, 2, 128), dtype=np.float32) for _ in range(2)]
    vs = [rng.standard_normal((1, 2, 128), dtype=np.float32) for _ in range(2)]
    got = run_gpu(torch_cuda, pack_paged(q, ks, vs))
    for b in range(2):
        vb = W.bf16_bits_to_f64(W.f32_to_bf16_bits(vs[b]))[0]
        for h in range(8):
            assert np.array_equal(got[b, h].astype(np.float64), vb[h // 4])
    for L in (17, 33, 250):
        q0 = np.zeros((1, 4, 64), dtype=np.float32)
        k = [rng.standard_normal((L, 1, 64), dtype=np.float32)]
        v = [rng.integers(-8, 8, size=(L, 1, 64), endpoint=True).astype(np.float32)]
        got = run_gpu(torch_cuda, pack_paged(q0, k, v))
        assert np.abs(got[0, 0] - v[0].astype(np.float64).mean(axis=0)[0]).max() < 1e-5


def test_determinism_and_page_permutation(torch_cuda):
    rng = np.random.default_rng(5)
    lens = [300, 17, 2000, 64]
    q = rng.standard_normal((4, 8, 64), dtype=np.float32)
    ks = [rng.standard_normal((L, 2, 64), dtype=np.float32) for L in lens]
    vs = [rng.standard_normal((L, 2, 64), dtype=np.float32) for L in lens]
    a1, a2 = run_gpu(torch_cuda, pack_paged(q, ks, vs, seed=0, permute=False), repeat=2)
    assert np.array_equal(a1.view(np.uint32), a2.view(np.uint32))
    b = run_gpu(torch_cuda, pack_paged(q, ks, vs, seed=3, permute=True, slack=9))
    # same lengths -> same partition -> same arithmetic order: physical placement must not matter at all
    assert np.array_equal(a1.view(np.uint32), b.view(np.uint32))


def test_cu_budget_changes_split_not_result(torch_cuda, jo):
    w = W.build(W.SHAPES[3], [5000, 9000, 123], seed=2, cfg=91)
    ref = jo.decode_attention(*arrays(w))
    for budget in (1, 7, 64):
        check(run_gpu(torch_cuda, arrays(w), cu_budget=budget), ref, f"cu_budget {budget}")


@pytest.mark.parametrize("hq,hkv,d", [(32, 8, 128), (14, 2, 64), (5, 5, 64), (16, 1, 128)])   # wave groups of 8, 2, 1, 1
def test_two_level_merge_at_many_splits(torch_cuda, jo, hq, hkv, d):
    # sequences cut into 16 pieces or more are merged cluster by cluster (8 wave groups each) and then over the
    # clusters; the CU budget moves the span, hence where the pieces, the cluster borders and the 16-piece limit fall:
    # long sequences that begin and end at every kind of place, short ones in between, twice on one handle
    lens = np.array([40000, 3, 25000, 100, 0, 17000, 17, 9000], dtype=np.int32)
    w = W.build(W.Shape("t", 0, hq, hkv, d, 1), lens, seed=31, cfg=93)
    ref = jo.decode_attention(*arrays(w))
    for budget in (0, 37, 64, 101, 160, 256):
        outs = run_gpu(torch_cuda, arrays(w), cu_budget=budget, repeat=2)
        check(outs[0], ref, f"two-level merge {hq}/{hkv}/{d} budget {budget}")
        assert np.array_equal(outs[0].view(np.uint32), outs[1].view(np.uint32)), f"budget {budget}: second call differs"


def walk_partition(lens, hkv, maxp, hdr, wave_start):
    """Walk every wave's share of the work line from where the library says it starts, in the documented line
    order (request-major over the requests that own pages, then kv-head group, then page; member i of a group of
    `wg` waves serves the kv heads i, i + wg, ...), and count how often each (request, kv head, page) is visited.
    Plain index work written for this test: it shares nothing with the library or with the oracle directory."""
    units, span, active, slots, wg = hdr[:5]
    n = np.minimum((np.asarray(lens, dtype=np.int64) + 15) // 16, maxp)
    n[np.asarray(lens) <= 0] = 0
    live = [int(b) for b in np.nonzero(n)[0]]
    nxt = {b: (live[i + 1] if i + 1 < len(live) else None) for i, b in enumerate(live)}
    seen = np.zeros((len(lens), hkv, max(1, int(n.max(initial=0)))), dtype=np.int32)
    owned = []
    for g in range(active):
        count = min(span, units - g * span)
        owned.append(count)
        for i in range(wg):
            b, kv, pg = wave_start[g * wg + i][:3]
            assert kv % wg == i and n[b] > 0 and 0 <= pg < n[b], (g, i, b, kv, pg)
            left = count
            while left > 0:
                take = min(left, int(n[b]) - pg)
                seen[b, kv, pg:pg + take] += 1
                left -= take
                pg += take
                if pg == n[b]:
                    pg, kv = 0, kv + wg
                    if kv >= hkv:
                        kv, b = i, nxt[b]
                        assert b is not None or left == 0, "a wave walked off the end of the work line"
    return n, seen, owned


@pytest.mark.parametrize("hkv,d", [(8, 128), (2, 64), (5, 64), (1, 128)])   # wave groups of 8 (4 on budgets that 8 does not divide), 2, 1 and 1
def test_partition_owns_every_page_exactly_once(torch_cuda, hkv, d):
    """The work partition pinned by validity on what the library itself returns: every (request, kv head, page)
    unit is owned by exactly one wave, every active group owns `span` units and the last one the remainder."""
    from paper_2604_23838_amd import binding as jb
    torch = torch_cuda
    rng = np.random.default_rng(3)
    shrinking = W.draw_seq_lens(2, np.random.default_rng(5)).copy()
    shrinking[rng.random(256) < 0.9] = 0                       # nine in ten requests have finished
    cases = [[17, 100, 250, 1000], [0, 0, 0], [1], [5, 0, 0, 70000, 3, 0], shrinking.tolist()]
    cases += [W.draw_seq_lens(cfg, np.random.default_rng(seed)).tolist() for cfg, seed in ((2, 0), (3, 0), (5, 0), (3, 2))]
    for lens in cases:
        B, maxp = len(lens), 2048                              # 70000 tokens exceed 16 * 2048: clamped and flagged
        for budget in (0, 3, 64):
            op = jb.DecodeAttention(B, hkv * 4, hkv, d, maxp, 64, cu_budget=budget)
            tl = torch.tensor(lens, dtype=torch.int32, device="cuda:0")
            hdr, ws, cum = op.partition(tl)
            units, span, active, slots, wg = hdr[:5]
            assert slots == jb.jd_wave_slots(op.handle) and slots % wg == 0
            want = 1                                           # the largest power of two up to 8 dividing heads and slots
            while want < 8 and hkv % (2 * want) == 0 and slots % (2 * want) == 0:
                want *= 2
            assert wg == want
            n, seen, owned = walk_partition(lens, hkv, maxp, hdr, ws)
            assert units == int(n.sum()) * (hkv // wg)
            assert cum == np.concatenate([[0], np.cumsum(n)]).tolist()
            assert active * wg <= slots and span >= 1
            assert active == (units + span - 1) // span
            assert all(c == span for c in owned[:-1]) and (not owned or 0 < owned[-1] <= span)
            for b in range(B):
                assert (seen[b, :, :n[b]] == 1).all(), f"request {b}: a page is owned {seen[b].max()} times or never"
                assert (seen[b, :, n[b]:] == 0).all()
            assert all(r == [0, 0, 0, 0] for r in ws[active * wg:])
            if max(lens) > maxp * 16:
                with pytest.raises(jb.JdError) as e:
                    op.check_flags()
                assert "sequence length" in str(e.value)
            op.close()


def test_bad_page_id_is_flagged_not_dereferenced(torch_cuda):
    from paper_2604_23838_amd import binding as jb
    w = W.gen_config(1, 0)
    bt = w.block_table.copy()
    bt[2, 3] = w.num_pages + 12345
    bt[1, 0] = -7
    with pytest.raises(jb.JdError) as e:
        run_gpu(torch_cuda, (w.q, w.k_pages, w.v_pages, bt, w.seq_lens))
    assert e.value.status == jb.JD_ERR_BAD_INPUT
    assert "block-table entry" in str(e.value)


def test_misaligned_and_null_arguments_are_refused_before_any_launch(torch_cuda):
    """Every refusal below happens on the host; the addresses are never handed to a kernel."""
    torch = torch_cuda
    from paper_2604_23838_amd import binding as jb
    cfg = jb.jd_config(batch=2, num_q_heads=4, num_kv_heads=2, head_dim=64, page_size=16, max_pages_per_seq=4,
                       num_pages=8, softmax_scale=0.0, cu_budget=0)
    h = jb.jd_create(cfg)
    try:
        buf = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
        a = buf.data_ptr()
        assert a % 16 == 0
        ok = dict(q=a, k=a + 4096, v=a + 8192, bt=a + 12288, sl=a + 16384, out=a + 20480, ql=a + 24576, qo=a + 28672)
        for bad in ("q", "k", "v", "out"):
            args = dict(ok); args[bad] += 8
            with pytest.raises(jb.JdError) as e:
                jb.jd_decode_attention(h, args["q"], args["k"], args["v"], args["bt"], args["sl"], args["out"])
            assert e.value.status == jb.JD_ERR_INVALID_ARG, bad
        for bad in ("bt", "sl"):
            args = dict(ok); args[bad] += 2
            with pytest.raises(jb.JdError) as e:
                jb.jd_decode_attention(h, args["q"], args["k"], args["v"], args["bt"], args["sl"], args["out"])
            assert e.value.status == jb.JD_ERR_INVALID_ARG, bad
        for bad in ("bt", "sl", "ql", "qo"):
            args = dict(ok); args[bad] += 2
            with pytest.raises(jb.JdError) as e:
                jb.jd_prefill_attention(h, args["q"], args["k"], args["v"], args["bt"], args["sl"], args["ql"],
                                        args["qo"], 16, 16, args["out"])
            assert e.value.status == jb.JD_ERR_INVALID_ARG, bad
        with pytest.raises(jb.JdError) as e:
            jb.jd_append_kv(h, ok["q"], ok["q"], ok["k"], ok["v"], ok["bt"], ok["sl"] + 2)
        assert e.value.status == jb.JD_ERR_INVALID_ARG
        with pytest.raises(jb.JdError) as e:
            jb.jd_decode_attention(h, ok["q"], None, ok["v"], ok["bt"], ok["sl"], ok["out"])
        assert e.value.status == jb.JD_ERR_INVALID_ARG
        assert "non-NULL" in str(e.value)
    finally:
        jb.jd_destroy(h)


def test_random_shapes(torch_cuda, jo):
    # a seeded sweep over head layouts, group sizes up to 16, both head sizes and mixed length patterns
    rng = np.random.default_rng(2024)
    heads = [(1, 1), (2, 1), (3, 1), (5, 5), (6, 2), (8, 8), (12, 4), (16, 2), (16, 1), (24, 8), (40, 8), (48, 16), (64, 4)]
    for case in range(36):
        Hq, Hkv = heads[rng.integers(len(heads))]
        D = int(rng.choice([64, 128]))
        B = int(rng.integers(1, 40))
        kind = case % 4
        if kind == 0:
            lens = rng.integers(0, 40, size=B)
        elif kind == 1:
            lens = np.floor(rng.lognormal(np.log(300.0), 1.5, size=B)).clip(0, 12000)
        elif kind == 2:
            lens = rng.choice([0, 1, 15, 16, 17, 255, 256, 257, 4095], size=B)
        else:
            lens = np.where(rng.random(B) < 0.8, 0, rng.integers(1, 6000, size=B))
        lens = lens.astype(np.int32)
        shp = W.Shape(f"rand{case}", B, Hq, Hkv, D, 1)
        w = W.build(shp, lens, seed=case, cfg=200 + case)
        ref = jo.decode_attention(*arrays(w))
        budget = int(rng.choice([0, 0, 2, 33]))
        print(f"case {case}: B={B} Hq={Hq} Hkv={Hkv} D={D} kind={kind} budget={budget}", flush=True)
        check(run_gpu(torch_cuda, arrays(w), cu_budget=budget), ref, f"random case {case}")


def test_handle_reuse_with_changing_lengths(torch_cuda, jo):
    # one handle, one pool, three steps whose lengths (hence partition, split sequences and partial records)
    # differ: records and arrival counters left by one call must not leak into the next
    from paper_2604_23838_amd import binding as jb
    torch = torch_cuda
    shp = W.SHAPES[2]
    w = W.build(shp, [9000, 40, 3000, 700, 16, 5000, 1, 260], seed=4, cfg=92)
    tq, tk, tv, tbt, tl = to_dev(torch, arrays(w))
    op = jb.DecodeAttention(8, shp.num_q_heads, shp.num_kv_heads, shp.head_dim, w.max_pages_per_seq, w.num_pages)
    rng = np.random.default_rng(0)
    for step in range(4):
        lens = w.seq_lens.copy() if step == 0 else np.minimum(w.seq_lens, rng.integers(0, 9001, size=8)).astype(np.int32)
        if step == 2:
            lens[:] = [0, 0, 2999, 0, 0, 0, 1, 0]
        tl.copy_(torch.from_numpy(lens))
        out = torch.full((8, shp.num_q_heads, shp.head_dim), float("nan"), dtype=torch.float32, device="cuda:0")
        op(tq, tk, tv, tbt, tl, out)
        torch.cuda.synchronize()
        ref = jo.decode_attention(w.q, w.k_pages, w.v_pages, w.block_table, lens)
        check(out.cpu().numpy(), ref, f"reuse step {step}")
    op.check_flags()
    op.close()


def test_hip_graph_capture_and_replay(torch_cuda, jo):
    # the call only enqueues kernels, so it can be captured; every replay (with the program's own eager work and
    # synchronisations in between, and with new lengths written into the captured buffers) must match the oracle
    from paper_2604_23838_amd import binding as jb
    torch = torch_cuda
    shp = W.SHAPES[5]
    w = W.build(shp, [300, 2500, 17, 64, 1200, 8000], seed=6, cfg=93)
    tq, tk, tv, tbt, tl = to_dev(torch, arrays(w))
    B = 6
    op = jb.DecodeAttention(B, shp.num_q_heads, shp.num_kv_heads, shp.head_dim, w.max_pages_per_seq, w.num_pages)
    out = torch.zeros((B, shp.num_q_heads, shp.head_dim), dtype=torch.float32, device="cuda:0")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        op(tq, tk, tv, tbt, tl, out)      # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    eager = out.cpu().numpy().copy()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        op(tq, tk, tv, tbt, tl, out)
    rng = np.random.default_rng(1)
    lens = w.seq_lens.copy()
    for rep in range(4):
        if rep:
            lens = np.minimum(w.seq_lens, rng.integers(1, 8001, size=B)).astype(np.int32)
            tl.copy_(torch.from_numpy(lens))
        out.fill_(float("nan"))          # eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        ref = jo.decode_attention(w.q, w.k_pages, w.v_pages, w.block_table, lens)
        check(got, ref, f"graph replay {rep}")
        if rep == 0:
            assert np.array_equal(got.view(np.uint32), eager.view(np.uint32))
    op.check_flags()
    op.close()


FULL = {2: "qwen3-8b-like", 3: "stragglers", 4: "qwen3-32b-like", 5: "qwen2.5-0.5b-like"}


@pytest.mark.parametrize("cfg,seed", [(c, 0) for c in sorted(FULL)] + [(2, 1), (3, 2), (4, 1), (5, 1)])
def test_full_size_configs(torch_cuda, jo, cfg, seed):
    # the benchmark's workloads at full size, in the launch configuration bench.py times;
    # seed 0 is the headline draw, the others are the generator's further draws of lengths and pages
    w = W.gen_config(cfg, seed)
    got = run_gpu(torch_cuda, arrays(w))
    ref = jo.decode_attention(*arrays(w))
    check(got, ref, f"cfg{cfg} {FULL[cfg]} seed {seed}")


@pytest.mark.parametrize("n", [2, 4, 8])
def test_merged_straggler_batches(torch_cuda, jo, n):
    # Long-tail migration aggregates the stragglers of n data-parallel workers on one target (Sub-stage Merging):
    # the benchmark's merged batches at full size (n straggler draws of 8 requests x 16-32 k tokens in one batch,
    # up to 1.6 M tokens), checked against the oracle on sampled output rows: every request's first and last
    # query head and random ones in between
    lens = np.concatenate([W.draw_seq_lens(3, np.random.default_rng(i)) for i in range(n)])
    shp = W.SHAPES[3]
    w = W.build(W.Shape(f"merged{n}", len(lens), shp.num_q_heads, shp.num_kv_heads, shp.head_dim, 1), lens, seed=0,
                cfg=30 + n, threads=16)
    got = run_gpu(torch_cuda, arrays(w))
    rng = np.random.default_rng(40 + n)
    rows = [(b, h) for b in range(len(lens)) for h in (0, shp.num_q_heads - 1, *rng.integers(0, shp.num_q_heads, size=2))]
    rows = np.array(rows, dtype=np.int32)
    ref = jo.decode_attention(*arrays(w), rows=rows)
    check(got[rows[:, 0], rows[:, 1]], ref, f"merged stragglers n={n} ({len(rows)} sampled rows of {w.total_tokens} tokens)")


@pytest.mark.parametrize("hq,hkv,d", [(14, 2, 64), (16, 1, 64), (32, 8, 128)])
def test_closed_forms_on_long_sequences(torch_cuda, hq, hkv, d):
    # Closed forms where the steady loop does the work (with 64-wide heads: pairs of pages consumed as one softmax
    # update).  A zero query gives the mean of V over exactly L tokens (integer-valued V, so the mean is known to
    # fp32 rounding); one key that dominates all others, sitting in the middle of the sequence, returns its V row
    # exactly, wherever the running maximum was before it arrived.
    rng = np.random.default_rng(77)
    for L in (511, 512, 513, 4097):
        q0 = np.zeros((1, hq, d), dtype=np.float32)
        k = [rng.standard_normal((L, hkv, d), dtype=np.float32)]
        v = [rng.integers(-8, 8, size=(L, hkv, d), endpoint=True).astype(np.float32)]
        got = run_gpu(torch_cuda, pack_paged(q0, k, v, seed=L))
        want = v[0].astype(np.float64).mean(axis=0)                      # [hkv, d]
        for h in range(hq):
            assert np.abs(got[0, h] - want[h // (hq // hkv)]).max() < 2e-5, (L, h)
    L, hot = 3000, 1717
    q = np.zeros((1, hq, d), dtype=np.float32)
    q[:, :, 0] = 64.0
    k = rng.standard_normal((L, hkv, d)).astype(np.float32) * 0.25
    k[:, :, 0] = 0.0
    k[hot, :, 0] = 64.0                                                 # score 4096 * scale against ~0 elsewhere
    v = rng.standard_normal((L, hkv, d), dtype=np.float32)
    got = run_gpu(torch_cuda, pack_paged(q, [k], [v], seed=5))
    vb = W.bf16_bits_to_f64(W.f32_to_bf16_bits(v))[hot]
    for h in range(hq):
        assert np.array_equal(got[0, h].astype(np.float64), vb[h // (hq // hkv)]), h
