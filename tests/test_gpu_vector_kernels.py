"""GPU parity of the vector-ALU comparison kernels (jd_bench_decode_attention_vector) against the fp64 oracle.

These kernels are the path the matrix-core kernel was measured against; they are kept runnable for that
comparison and are not part of the product call.  Same tolerance as the product path.
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
    check(run_gpu(torch_cuda, arrays(w), vector_kernels=True), jo.decode_attention(*arrays(w)), "cfg1 vector")


@pytest.mark.parametrize("shape", [(8, 2, 64), (14, 2, 64), (32, 8, 128), (64, 8, 128), (4, 4, 128)])
def test_edge_lengths(torch_cuda, jo, shape):
    Hq, Hkv, D = shape
    edge = [[1], [15], [16], [17], [31, 32, 33], [0, 5, 0], [0, 0, 0], [1000, 1, 0, 64, 65], [63, 0, 0, 0, 0, 0, 0, 2049]]
    for i, lens in enumerate(edge):
        rng = np.random.default_rng(1000 + i)
        q = rng.standard_normal((len(lens), Hq, D), dtype=np.float32)
        ks = [rng.standard_normal((L, Hkv, D), dtype=np.float32) for L in lens]
        vs = [rng.standard_normal((L, Hkv, D), dtype=np.float32) for L in lens]
        arrs = pack_paged(q, ks, vs, seed=i)
        check(run_gpu(torch_cuda, arrs, vector_kernels=True), jo.decode_attention(*arrs), f"edge {lens} {shape} vector")


def test_group_size_outside_the_set_is_refused(torch_cuda):
    from paper_2604_23838_amd import binding as jb
    w = W.build(W.Shape("g3", 0, 6, 2, 64, 1), [40, 3], seed=1, cfg=95)
    with pytest.raises(jb.JdError) as e:
        run_gpu(torch_cuda, arrays(w), vector_kernels=True)
    assert e.value.status == jb.JD_ERR_UNSUPPORTED


def test_ragged_batch_and_both_paths_on_one_handle(torch_cuda, jo):
    # long-tailed lengths spanning many spans; the product call and the comparison kernels alternate on one
    # handle (separate tables, one flag word), with lengths that change in between
    from paper_2604_23838_amd import binding as jb
    torch = torch_cuda
    rng = np.random.default_rng(7)
    lens = np.clip(np.floor(rng.lognormal(np.log(600.0), 1.3, size=96)), 1, 20000).astype(np.int32)
    lens[5] = 0
    for shp in (W.SHAPES[2], W.SHAPES[5]):
        w = W.build(shp, lens, seed=7, cfg=90)
        tq, tk, tv, tbt, tl = to_dev(torch, arrays(w))
        op = jb.DecodeAttention(len(lens), shp.num_q_heads, shp.num_kv_heads, shp.head_dim, w.max_pages_per_seq, w.num_pages)
        for step, vec in enumerate((True, False, True, False)):
            cur = lens if step < 2 else np.minimum(lens, rng.integers(0, 3000, size=len(lens))).astype(np.int32)
            tl.copy_(torch.from_numpy(cur))
            out = torch.full((len(lens), shp.num_q_heads, shp.head_dim), float("nan"), dtype=torch.float32, device="cuda:0")
            op(tq, tk, tv, tbt, tl, out, vector_kernels=vec)
            torch.cuda.synchronize()
            ref = jo.decode_attention(w.q, w.k_pages, w.v_pages, w.block_table, cur)
            check(out.cpu().numpy(), ref, f"ragged {shp.name} step {step} {'vector' if vec else 'product'}")
        op.check_flags()
        op.close()


def test_bad_page_id_is_flagged(torch_cuda):
    from paper_2604_23838_amd import binding as jb
    w = W.gen_config(1, 0)
    bt = w.block_table.copy()
    bt[2, 3] = w.num_pages + 12345
    with pytest.raises(jb.JdError) as e:
        run_gpu(torch_cuda, (w.q, w.k_pages, w.v_pages, bt, w.seq_lens), vector_kernels=True)
    assert e.value.status == jb.JD_ERR_BAD_INPUT


@pytest.mark.parametrize("cfg", [3, 5])
def test_full_size_configs(torch_cuda, jo, cfg):
    w = W.gen_config(cfg, 0)
    check(run_gpu(torch_cuda, arrays(w), vector_kernels=True), jo.decode_attention(*arrays(w)), f"cfg{cfg} vector")
