"""CU-budgeted decode on a stream that is itself confined to a subset of the compute units.

The paper runs co-located sub-stages in SM partitions and replays one pre-recorded graph per SM budget
(Sub-stage Multiplexing, "Dynamic Resource Allocation").  Here: a stream with a CU mask of 25 / 50 / 75 % of
the device, a handle whose cu_budget is the mask's CU count (one workgroup per unit of the partition), the
straggler batch and a rollout-shaped batch, eagerly and as a replayed HIP graph, against the oracle.
"""
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


def test_mask_sizes_outside_the_set_are_refused(torch_cuda):
    from paper_2604_23838_amd import binding as jb
    for n in (0, 8, 100, 1 << 20):
        with pytest.raises(jb.JdError) as e:
            jb.jd_bench_stream_create_cu_masked(n)
        assert e.value.status == jb.JD_ERR_INVALID_ARG


@pytest.mark.parametrize("pct", [25, 50, 75])
def test_decode_on_a_cu_masked_stream(torch_cuda, jo, pct):
    from paper_2604_23838_amd import binding as jb
    torch = torch_cuda
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    n_cus = cus * pct // 100
    handle = jb.jd_bench_stream_create_cu_masked(n_cus)
    stream = torch.cuda.ExternalStream(handle)
    rng = np.random.default_rng(pct)
    rollout = (512 + np.minimum(np.floor(rng.lognormal(np.log(2048.0), 1.0, size=48)), 16384)).astype(np.int32)
    workloads = [("stragglers", W.gen_config(3, 0, threads=16)),
                 ("rollout-shaped", W.build(W.SHAPES[2], rollout, seed=pct, cfg=97, threads=16))]
    try:
        for name, w in workloads:
            s = w.shape
            t = to_dev(torch, arrays(w))
            ref = jo.decode_attention(*arrays(w))
            op = jb.DecodeAttention(s.batch, s.num_q_heads, s.num_kv_heads, s.head_dim, w.max_pages_per_seq, w.num_pages,
                                    cu_budget=n_cus)
            assert jb.jd_wave_slots(op.handle) == 4 * n_cus
            out = torch.full((s.batch, s.num_q_heads, s.head_dim), float("nan"), dtype=torch.float32, device="cuda:0")
            torch.cuda.synchronize()
            with torch.cuda.stream(stream):
                op(*t, out)                       # eager, on the confined stream
            stream.synchronize()
            eager = out.cpu().numpy().copy()
            check(eager, ref, f"{name} eager on {n_cus} of {cus} CUs")
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                op(*t, out)
            lens = w.seq_lens.copy()
            for rep in range(3):
                if rep:                           # new lengths in the captured buffer, eager work in between
                    lens = np.maximum(1, w.seq_lens - rng.integers(0, 4000, size=s.batch)).astype(np.int32)
                    t[4].copy_(torch.from_numpy(lens))
                out.fill_(float("nan"))
                torch.cuda.synchronize()
                with torch.cuda.stream(stream):
                    g.replay()
                stream.synchronize()
                torch.cuda.synchronize()
                got = out.cpu().numpy()
                check(got, jo.decode_attention(w.q, w.k_pages, w.v_pages, w.block_table, lens),
                      f"{name} graph replay {rep} on {n_cus} CUs")
                if rep == 0:
                    assert np.array_equal(got.view(np.uint32), eager.view(np.uint32))
            del g
            op.check_flags(stream)
            op.close()
    finally:
        torch.cuda.synchronize()
        jb.jd_bench_stream_destroy(handle)


def test_grid_larger_than_the_partition_runs_in_two_passes(torch_cuda, jo):
    # A handle sized for 128 units on a stream confined to 64: the second half of the workgroups only starts when
    # the first half has finished.  Nothing in the kernel waits for another workgroup, so the step completes; and the
    # pieces that second-pass waves announce early are then the last of their streams to be counted, which is the
    # path on which the announcing wave itself has to find that out at its end and merge.
    from paper_2604_23838_amd import binding as jb
    torch = torch_cuda
    handle = jb.jd_bench_stream_create_cu_masked(64)
    stream = torch.cuda.ExternalStream(handle)
    try:
        for w in (W.gen_config(3, 1, threads=16), W.build(W.SHAPES[5], W.draw_seq_lens(5, np.random.default_rng(4))[:300],
                                                          seed=4, cfg=97, threads=16)):
            s = w.shape
            t = to_dev(torch, arrays(w))
            ref = jo.decode_attention(*arrays(w))
            op = jb.DecodeAttention(s.batch, s.num_q_heads, s.num_kv_heads, s.head_dim, w.max_pages_per_seq, w.num_pages,
                                    cu_budget=128)
            out = torch.full((s.batch, s.num_q_heads, s.head_dim), float("nan"), dtype=torch.float32, device="cuda:0")
            torch.cuda.synchronize()
            for rep in range(2):
                with torch.cuda.stream(stream):
                    op(*t, out)
                stream.synchronize()
                check(out.cpu().numpy(), ref, f"{s.name}: 128 workgroups on 64 units, call {rep}")
                out.fill_(float("nan"))
                torch.cuda.synchronize()
            op.check_flags(stream)
            op.close()
    finally:
        torch.cuda.synchronize()
        jb.jd_bench_stream_destroy(handle)
