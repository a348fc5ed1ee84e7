"""The allocation-free entry point jd_decode_attention_static against jd_decode_attention on a handle (same
kernels, other workspace: bitwise the same result) and against the oracle, on two calls in a row, the second
with a smaller input, so that whatever the static array kept from the first call must not show."""
import numpy as np
import pytest

from paper_2604_23838_amd import workloads as W
from gpu_helpers import arrays, check, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (run with -m 'not gpu' elsewhere)")
    return torch


def both_ways(torch, jb, w):
    s = w.shape
    t = to_dev(torch, arrays(w))
    cfg = jb.jd_config(s.batch, s.num_q_heads, s.num_kv_heads, s.head_dim, 16, w.max_pages_per_seq, w.num_pages, 0.0, 0)
    out_static = torch.full((s.batch, s.num_q_heads, s.head_dim), float("nan"), dtype=torch.float32, device="cuda:0")
    out_handle = torch.full_like(out_static, float("nan"))
    stream = torch.cuda.current_stream().cuda_stream
    jb.jd_decode_attention_static(cfg, t[0].data_ptr(), t[1].data_ptr(), t[2].data_ptr(), t[3].data_ptr(),
                                  t[4].data_ptr(), out_static.data_ptr(), stream)
    torch.cuda.synchronize()
    op = jb.DecodeAttention(s.batch, s.num_q_heads, s.num_kv_heads, s.head_dim, w.max_pages_per_seq, w.num_pages)
    op(*t, out_handle)
    torch.cuda.synchronize()
    op.check_flags()
    op.close()
    return out_static.cpu().numpy(), out_handle.cpu().numpy()


def test_static_entry_point_matches_the_handle_twice(torch_cuda, jo):
    from paper_2604_23838_amd import binding as jb
    torch = torch_cuda
    rng = np.random.default_rng(31)
    # first call: long sequences cut into many pieces (records and arrival counters in use all over the array);
    # second call: a smaller batch of another head shape, shorter, with an empty request and split sequences again
    big = W.build(W.SHAPES[2], np.array([9000, 40, 3000, 700, 16, 5000, 1, 260, 12000, 77, 2049, 6000], dtype=np.int32),
                  seed=31, cfg=98)
    small = W.build(W.SHAPES[5], np.array([1500, 0, 33, 4000, 17], dtype=np.int32), seed=32, cfg=98)
    for name, w in (("first (larger) call", big), ("second (smaller) call", small)):
        got_static, got_handle = both_ways(torch, jb, w)
        ref = jo.decode_attention(*arrays(w))
        check(got_static, ref, f"static entry point, {name}")
        check(got_handle, ref, f"handle, {name}")
        assert np.array_equal(got_static.view(np.uint32), got_handle.view(np.uint32)), name


def test_static_entry_point_under_graph_capture(torch_cuda, jo):
    # the callers this entry point is for: captured once (after a first call outside the capture has resolved the
    # array's address), replayed with the program's own eager work in between and new lengths in the captured buffer
    from paper_2604_23838_amd import binding as jb
    torch = torch_cuda
    w = W.build(W.SHAPES[5], np.array([300, 2500, 17, 64, 1200, 8000], dtype=np.int32), seed=6, cfg=93)
    s = w.shape
    t = to_dev(torch, arrays(w))
    cfg = jb.jd_config(s.batch, s.num_q_heads, s.num_kv_heads, s.head_dim, 16, w.max_pages_per_seq, w.num_pages, 0.0, 0)
    out = torch.zeros((s.batch, s.num_q_heads, s.head_dim), dtype=torch.float32, device="cuda:0")

    def call():
        jb.jd_decode_attention_static(cfg, t[0].data_ptr(), t[1].data_ptr(), t[2].data_ptr(), t[3].data_ptr(),
                                      t[4].data_ptr(), out.data_ptr(), torch.cuda.current_stream().cuda_stream)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        call()
    rng = np.random.default_rng(2)
    lens = w.seq_lens.copy()
    for rep in range(4):
        if rep:
            lens = np.minimum(w.seq_lens, rng.integers(1, 8001, size=s.batch)).astype(np.int32)
            t[4].copy_(torch.from_numpy(lens))
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        check(out.cpu().numpy(), jo.decode_attention(w.q, w.k_pages, w.v_pages, w.block_table, lens), f"static entry point, replay {rep}")


def test_static_entry_point_rejects_what_does_not_fit(torch_cuda):
    from paper_2604_23838_amd import binding as jb
    torch = torch_cuda
    buf = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    a = buf.data_ptr()
    # group size 16 with 128-wide heads on the library's default share of the compute units: 2 records of
    # 16 x 130 floats per wave slot exceed the 12 MiB array
    cfg = jb.jd_config(4, 64, 4, 128, 16, 8, 64, 0.0, 0)
    with pytest.raises(jb.JdError) as e:
        jb.jd_decode_attention_static(cfg, a, a + 4096, a + 8192, a + 12288, a + 16384, a + 20480)
    assert e.value.status == jb.JD_ERR_UNSUPPORTED and "static array holds" in str(e.value)
    cfg.head_dim = 96
    with pytest.raises(jb.JdError) as e:
        jb.jd_decode_attention_static(cfg, a, a + 4096, a + 8192, a + 12288, a + 16384, a + 20480)
    assert e.value.status == jb.JD_ERR_UNSUPPORTED
    cfg = jb.jd_config(4, 8, 2, 64, 16, 8, 64, 0.0, 0)
    with pytest.raises(jb.JdError) as e:
        jb.jd_decode_attention_static(cfg, a + 8, a + 4096, a + 8192, a + 12288, a + 16384, a + 20480)
    assert e.value.status == jb.JD_ERR_INVALID_ARG
