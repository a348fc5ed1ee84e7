"""GPU parity of jd_append_kv (byte work: bit-exact against the plain-Python reference) and of the closed
decode loop append -> attention against the fp64 oracle."""
import numpy as np
import pytest

from oracle import append_ref
from paper_2604_23838_amd import workloads as W
from helpers import error_report

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    return torch


def bf16_dev(torch, a):
    return torch.from_numpy(a.view(np.int16)).to("cuda:0").view(torch.bfloat16)


def bits_host(torch, t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def token_rows(w, lens):
    """K and V rows ([B, Hkv, D] bit patterns) of token position lens[b] of every request (zeros where the
    request has no such token in the generated pool)."""
    s = w.shape
    k = np.zeros((s.batch, s.num_kv_heads, s.head_dim), dtype=np.uint16)
    v = np.zeros_like(k)
    for b in range(s.batch):
        L = int(lens[b])
        if L < int(w.seq_lens[b]):
            pg = int(w.block_table[b, L // 16])
            k[b] = w.k_pages[pg, :, L % 16, :]
            v[b] = w.v_pages[pg, :, L % 16, :]
    return k, v


@pytest.mark.parametrize("shape_id", [2, 5])
def test_closed_decode_loop(torch_cuda, jo, shape_id):
    # Start every request T tokens short of its generated length with those tokens wiped from the pool, then
    # decode T steps: each step appends the original rows back and attends.  The pool and the lengths must
    # follow the reference bit for bit, the attention output the oracle; at the end the pool is the original.
    from paper_2604_23838_amd import binding as jb
    torch = torch_cuda
    shp = W.SHAPES[shape_id]
    full = np.array([40, 16, 333, 1, 2049, 700, 32, 17], dtype=np.int32)
    w = W.build(shp, full, seed=21, cfg=95, poison=True)
    T = 18
    start = np.maximum(full - T, 0).astype(np.int32)
    start[3] = 0                      # a finished slot: never appended to without a mask
    kp, vp = w.k_pages.copy(), w.v_pages.copy()
    for b in range(len(full)):        # wipe what will be appended
        for j in range(int(start[b]), int(full[b])):
            pg = int(w.block_table[b, j // 16])
            kp[pg, :, j % 16, :] = W.BF16_NAN
            vp[pg, :, j % 16, :] = W.BF16_NAN
    B = len(full)
    tq, tk, tv = bf16_dev(torch, w.q), bf16_dev(torch, kp), bf16_dev(torch, vp)
    tbt = torch.from_numpy(w.block_table).to("cuda:0")
    tl = torch.from_numpy(start).to("cuda:0")
    op = jb.DecodeAttention(B, shp.num_q_heads, shp.num_kv_heads, shp.head_dim, w.max_pages_per_seq, w.num_pages)
    ref_k, ref_v, ref_l = kp, vp, start
    for step in range(T):
        kn, vn = token_rows(w, ref_l)
        # a request that has reached its generated length stops.  While none has, alternate between the explicit
        # mask and the NULL-mask rule (append wherever L > 0); afterwards the mask is needed.
        running = ((ref_l < full) & (ref_l > 0)).astype(np.int32)
        nobody_done = bool(((ref_l < full) | (ref_l == 0)).all())
        use_mask = (step % 2 == 1) or not nobody_done
        active = running if use_mask else None
        tact = torch.from_numpy(running).to("cuda:0") if use_mask else None
        op.append(bf16_dev(torch, kn), bf16_dev(torch, vn), tk, tv, tbt, tl, tact)
        ref_k, ref_v, ref_l = append_ref.append_kv(kn, vn, ref_k, ref_v, w.block_table, ref_l, active)
        out = op(tq, tk, tv, tbt, tl)
        torch.cuda.synchronize()
        assert np.array_equal(tl.cpu().numpy(), ref_l), f"lengths differ at step {step}"
        ref = jo.decode_attention(w.q, ref_k, ref_v, w.block_table, ref_l)
        ma, mr = error_report(out.cpu().numpy(), ref)
        assert np.isfinite(out.cpu().numpy()).all() and ma <= 5e-3 and mr <= 1e-2, (step, ma, mr)
    assert np.array_equal(bits_host(torch, tk), ref_k) and np.array_equal(bits_host(torch, tv), ref_v)
    grown = np.where(start > 0, full, 0)   # slots that started empty are finished rows and stay empty
    assert np.array_equal(ref_l, grown) and (grown > 0).sum() >= 5
    # every appended slot carries its original bits again
    for b in range(B):
        for j in range(int(start[b]), int(grown[b])):
            pg = int(w.block_table[b, j // 16])
            assert np.array_equal(ref_k[pg, :, j % 16, :], w.k_pages[pg, :, j % 16, :])
    op.check_flags()
    op.close()


def test_append_at_capacity_and_bad_page_are_flagged(torch_cuda):
    from paper_2604_23838_amd import binding as jb
    torch = torch_cuda
    shp = W.SHAPES[1]
    w = W.build(shp, [32, 5, 16], seed=3, cfg=96, poison=False)   # MAXP = 2: request 0 is full
    bt = w.block_table.copy()
    bt[2, 1] = w.num_pages + 7                                     # request 2 appends into an unassigned page
    tk, tv = bf16_dev(torch, w.k_pages), bf16_dev(torch, w.v_pages)
    tbt = torch.from_numpy(bt).to("cuda:0")
    tl = torch.from_numpy(w.seq_lens.copy()).to("cuda:0")
    rng = np.random.default_rng(0)
    kn = W.f32_to_bf16_bits(rng.standard_normal((3, shp.num_kv_heads, shp.head_dim), dtype=np.float32))
    vn = W.f32_to_bf16_bits(rng.standard_normal((3, shp.num_kv_heads, shp.head_dim), dtype=np.float32))
    op = jb.DecodeAttention(3, shp.num_q_heads, shp.num_kv_heads, shp.head_dim, 2, w.num_pages)
    op.append(bf16_dev(torch, kn), bf16_dev(torch, vn), tk, tv, tbt, tl)
    torch.cuda.synchronize()
    rk, rv, rl = append_ref.append_kv(kn, vn, w.k_pages, w.v_pages, bt, w.seq_lens)
    assert rl.tolist() == [32, 6, 16]
    assert np.array_equal(tl.cpu().numpy(), rl)
    assert np.array_equal(bits_host(torch, tk), rk) and np.array_equal(bits_host(torch, tv), rv)
    with pytest.raises(jb.JdError) as e:
        op.check_flags()
    assert e.value.status == jb.JD_ERR_BAD_INPUT
    op.close()


def test_decode_loop_under_one_graph(torch_cuda, jo):
    # append + attention captured once and replayed: each replay advances every request by one token
    from paper_2604_23838_amd import binding as jb
    torch = torch_cuda
    shp = W.SHAPES[2]
    full = np.array([300, 47, 1500, 16], dtype=np.int32)
    w = W.build(shp, full, seed=5, cfg=97, poison=False)
    T = 6
    lens = (full - T).astype(np.int32)
    B = len(full)
    tq, tk, tv = bf16_dev(torch, w.q), bf16_dev(torch, w.k_pages), bf16_dev(torch, w.v_pages)
    tbt = torch.from_numpy(w.block_table).to("cuda:0")
    tl = torch.from_numpy(lens).to("cuda:0")
    tkn = torch.zeros((B, shp.num_kv_heads, shp.head_dim), dtype=torch.bfloat16, device="cuda:0")
    tvn = torch.zeros_like(tkn)
    out = torch.zeros((B, shp.num_q_heads, shp.head_dim), dtype=torch.float32, device="cuda:0")
    op = jb.DecodeAttention(B, shp.num_q_heads, shp.num_kv_heads, shp.head_dim, w.max_pages_per_seq, w.num_pages)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        op(tq, tk, tv, tbt, tl, out)          # warm-up of the attention launch outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        op.append(tkn, tvn, tk, tv, tbt, tl)
        op(tq, tk, tv, tbt, tl, out)
    # the capture itself does not run the kernels: the lengths are still T short
    assert np.array_equal(tl.cpu().numpy(), lens)
    for step in range(T):
        kn, vn = token_rows(w, lens)          # the original rows: the pool stays what the generator made
        tkn.copy_(bf16_dev(torch, kn))
        tvn.copy_(bf16_dev(torch, vn))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        lens = lens + 1
        assert np.array_equal(tl.cpu().numpy(), lens)
        ref = jo.decode_attention(w.q, w.k_pages, w.v_pages, w.block_table, lens)
        ma, mr = error_report(out.cpu().numpy(), ref)
        assert ma <= 5e-3 and mr <= 1e-2, (step, ma, mr)
    assert np.array_equal(bits_host(torch, tk), w.k_pages)
    op.check_flags()
    op.close()
